/*
 * libpard -- batched end-to-end latency estimate, drop decision and survivor
 * compaction for queued inference-pipeline requests, on one AMD MI355X (gfx950).
 *
 * The method is PARD's proactive request dropping (EuroSys '26), Section 3.2-3.3,
 * posed on a snapshot of the queues:
 *   - a request's end-to-end latency is split into preceding, current and subsequent
 *     modules (Eq.(1)); every module contributes queueing + batch wait + execution
 *     (Eq.(2)); the estimate is their sum along a downstream path (Eq.(4)) and, for a
 *     DAG pipeline, the maximum over all downstream paths (Section 3.2, last paragraph);
 *   - queues are ordered by remaining latency budget, lowest first (LBF) or highest
 *     first (HBF) (Section 3.3); arrival order (FCFS) is the paper's ablation (Section 5.3);
 *   - a request is dropped when the estimate says it cannot finish within its SLO.
 *
 * Snapshot form of the per-stage term, with `a` requests ahead in a stage with batch
 * size B, W workers and batch-latency table lat[1..64] (integer microseconds):
 *     cost(a) = floor( ceil(a / B) * lat[B] / W )  +  lat[ min(B, a + 1) ]
 * In the request's own stage `a` is its 0-based queue position after ordering; in every
 * downstream stage `a` is that stage's whole queue length.  estimate = max over the
 * source-to-sink paths through the request's stage of the summed costs from its stage
 * to the sink.  drop = (min(now + estimate, INT32_MAX) > deadline).  The estimate
 * itself is reported clamped to INT32_MAX.  Ties in the queue order are broken by
 * ascending request index.  A stage id outside [0, S) is read as the nearest valid one.
 *
 * Conventions
 *   - C ABI.  Every function returns PARD_OK (0) or a negative pard_status; nothing
 *     throws or aborts.
 *   - "host" pointers are ordinary CPU memory, read only during the call.
 *     "device" pointers are HIP device memory owned by the caller; they must stay
 *     valid until the work queued on `stream` has completed.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  The two
 *     hot calls only enqueue kernels: they do not allocate, free or synchronise.
 *   - A plan changes only through pard_plan_set_modes.  It may be used from several
 *     streams at once, provided each concurrent call has its own workspace.  Two
 *     exceptions: the sampled variant of pard_sub_latency, which stages its draws in
 *     scratch memory the plan owns (see there), and pard_compact where it compacts the
 *     queues as one stream (see there): its workgroups wait for each other and need the
 *     device's compute units to themselves.
 */
#ifndef PARD_H_
#define PARD_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PARD_LAT_ENTRIES 64      /* batch-latency table entries per stage: b = 1..64      */
#define PARD_MAX_STAGES 64       /* S <= 64                                               */
#define PARD_MAX_PATHS_PER_DAG 1024
#define PARD_MAX_PATH_ENTRIES_PER_DAG 8192   /* sum of path lengths of one DAG            */
#define PARD_MAX_WORKERS 1048576 /* W <= 2^20                                             */
#define PARD_FUSED_SNAPSHOT_CAPACITY 8192    /* snapshots up to this size are processed by
                                                one workgroup entirely in on-chip memory  */

typedef enum {
    PARD_OK = 0,
    PARD_E_NULL = -1,            /* a required pointer is NULL                            */
    PARD_E_BAD_SHAPE = -2,       /* K < 1, S outside 1..64, n < 0 or too large            */
    PARD_E_BAD_BATCH = -3,       /* a batch size outside 1..64                            */
    PARD_E_BAD_WORKERS = -4,     /* a worker count outside 1..PARD_MAX_WORKERS            */
    PARD_E_BAD_LATENCY = -5,     /* a negative latency                                    */
    PARD_E_BAD_DAG = -6,         /* edge out of range, self loop, cycle, bad row_ptr      */
    PARD_E_TOO_MANY_PATHS = -7,  /* path expansion exceeds the per-DAG limits above       */
    PARD_E_WORKSPACE = -8,       /* workspace NULL, misaligned or too small               */
    PARD_E_HIP = -9,             /* a HIP runtime call failed                             */
    PARD_E_BAD_MODE = -10,       /* order mode not one of PARD_ORDER_*                    */
    PARD_E_UNSUPPORTED = -11,    /* shape or value range not supported (see the calls)    */
    PARD_E_SCRATCH = -12         /* the call needs more than PARD_STATIC_SCRATCH_BYTES of the
                                    library's built-in scratch buffer                      */
} pard_status;

enum { PARD_ORDER_LBF = 0,       /* ascending deadline  (low remaining budget first)      */
       PARD_ORDER_HBF = 1,       /* descending deadline (high remaining budget first)     */
       PARD_ORDER_FCFS = 2 };    /* ascending arrival                                     */

typedef struct pard_plan pard_plan_t;    /* opaque; owned by the library until destroyed  */

/*
 * Pipeline description (Section 4 "Implementation": a pipeline is a set of modules with
 * predecessor/successor lists; Section 3.2: profiled batch latencies, batch sizes).
 * All arrays are HOST memory, int32.  D = dag_shared ? 1 : num_snapshots descriptions
 * are stored back to back.  The successor lists of DAG d are
 * dag_col[base_d + dag_row_ptr[d*(S+1)+s] .. base_d + dag_row_ptr[d*(S+1)+s+1]) where
 * dag_row_ptr[d*(S+1)] == 0 and base_d is the sum of the previous DAGs' edge counts.
 */
typedef struct {
    int32_t num_snapshots;       /* K >= 1                                                */
    int32_t num_stages;          /* S in 1..64, the same for every snapshot               */
    int32_t dag_shared;          /* 1: one description for all snapshots, 0: one each     */
    const int32_t* dag_row_ptr;  /* [D*(S+1)]                                             */
    const int32_t* dag_col;      /* successor stage ids (may be NULL when there are none) */
    const int32_t* batch;        /* [D*S]     B in 1..64                                  */
    const int32_t* workers;      /* [D*S]     W in 1..PARD_MAX_WORKERS                    */
    const int32_t* lat_us;       /* [D*S*64]  lat_us[(d*S+s)*64 + b-1] >= 0, b = 1..64    */
    const int32_t* order_mode;   /* [D*S]     PARD_ORDER_*                                */
} pard_plan_desc_t;

/*
 * Host-only validation and DAG -> path expansion (the DAG sentence of Section 3.2: the
 * estimate is taken along each subsequent path).  Touches no GPU.  On success writes
 * the number of source-to-sink paths summed over all D DAGs and the longest path in
 * stages.  Either output pointer may be NULL.  Errors: every PARD_E_BAD_* code,
 * PARD_E_NULL, PARD_E_TOO_MANY_PATHS.
 */
int pard_plan_check(const pard_plan_desc_t* desc, int64_t* total_paths, int32_t* max_path_len);

/*
 * Validates `desc` as pard_plan_check does, expands every DAG into its path CSR,
 * precomputes the per-stage constants and copies everything to the current HIP device
 * (synchronous; this is the cold path).  *out receives the plan.  The descriptor's
 * arrays are copied; the caller keeps ownership of them.
 */
int pard_plan_create(pard_plan_t** out, const pard_plan_desc_t* desc);

/* Frees the plan's device and host memory.  NULL is accepted. */
int pard_plan_destroy(pard_plan_t* plan);

/* Path statistics of a created plan (same meaning as in pard_plan_check). */
int pard_plan_info(const pard_plan_t* plan, int64_t* total_paths, int32_t* max_path_len);

/*
 * Bytes of device workspace pard_estimate_drop and pard_compact need for up to
 * max_requests requests in total and up to max_snapshot_requests in any one snapshot
 * (pass max_requests when unknown).  The workspace must be 256-byte aligned.  Its first
 * 32-bit word accumulates status bits (bit 0: a snapshot was larger than promised and was
 * truncated; no other bit is in use: no kernel of this library waits for another workgroup);
 * the caller zero-fills the workspace once after allocating it and may copy the word back at
 * any time.
 */
int pard_workspace_bytes(const pard_plan_t* plan, int64_t max_requests,
                         int64_t max_snapshot_requests, int64_t* bytes);

/*
 * Steps of the path: per-(snapshot, stage) queue lengths, segmented stable ordering
 * of the queues, queue positions, per-request estimate with the maximum over paths,
 * drop decision (Section 3.2 Eq.(1),(2),(4); Section 3.3 for the ordering).
 *
 *   n                      total requests, 0 <= n < 2^30
 *   max_snapshot_requests  caller's upper bound on snap_ptr[u+1]-snap_ptr[u]; selects the
 *                          on-chip path when <= PARD_FUSED_SNAPSHOT_CAPACITY, and there the
 *                          size of the workgroup that takes a snapshot (a tight bound is
 *                          faster: 64, 128, 256, 512, 1024, 2048, 4096, 8192 are the steps; up to
 *                          128 a single wave sorts the snapshot in registers).  A snapshot
 *                          larger than the promised bound is truncated to the bound and
 *                          raises bit 0 of the status word (memory safe, results for that
 *                          snapshot unspecified).
 *   d_arrival, d_deadline, d_stage   device int32[n], request order.  d_arrival may be
 *                          NULL when no stage of the plan uses PARD_ORDER_FCFS.
 *   d_snap_ptr             device int32[K+1], non-decreasing, snap_ptr[0]=0, snap_ptr[K]=n;
 *                          the requests of snapshot u are [snap_ptr[u], snap_ptr[u+1])
 *   d_now                  device int32[K], current time of each snapshot
 *   d_est                  device out int32[n]  estimate, request order, clamped to INT32_MAX
 *   d_drop                 device out uint8[n]  1 = drop, request order
 *   d_order                device out int32[n]  queue order: sorted position -> request id
 *   d_seg_ptr              device out int32[K*S+1] offsets of queue (u,s) inside d_order
 *
 * Errors: PARD_E_NULL, PARD_E_BAD_SHAPE, PARD_E_WORKSPACE, PARD_E_UNSUPPORTED (large
 * snapshots for which the bits of max_snapshot_requests - 1 plus the bits of K*S - 1
 * exceed 32), PARD_E_HIP.
 * Contents of the request arrays are not validated on the host.
 */
int pard_estimate_drop(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                       const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                       const int32_t* d_snap_ptr, const int32_t* d_now,
                       int32_t* d_est, uint8_t* d_drop, int32_t* d_order, int32_t* d_seg_ptr,
                       void* d_workspace, int64_t workspace_bytes, void* stream);

/*
 * pard_estimate_drop for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * kernels are the ones pard_estimate_drop launches; their workspace is a buffer of
 * PARD_STATIC_SCRATCH_BYTES that is part of the library's device image (each GPU the library
 * runs on holds its own copy until the process ends).  The call allocates and frees nothing.
 *
 *   d_status               device out uint32[1], may be NULL: receives the status bits the buffer has
 *                          accumulated since they were last taken (meaning as for the workspace's
 *                          first word); copied on `stream` after the kernels, then cleared
 *   everything else        as for pard_estimate_drop
 *
 * Snapshots up to PARD_FUSED_SNAPSHOT_CAPACITY need a few bytes of the buffer, so any n is
 * served; larger snapshots need what pard_workspace_bytes reports, and the call returns
 * PARD_E_SCRATCH when that exceeds PARD_STATIC_SCRATCH_BYTES (about 1.5 million requests).
 * All calls on one GPU share that GPU's buffer: two such calls that overlap in time on one GPU
 * (different streams) race; calls on one stream are ordered and safe.  The first call on a
 * device looks up the buffer's address (no allocation); make it outside a stream capture.
 * Errors: as pard_estimate_drop, plus PARD_E_SCRATCH.
 */
#define PARD_STATIC_SCRATCH_BYTES (32 << 20)
int pard_estimate_drop_static(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                              const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                              const int32_t* d_snap_ptr, const int32_t* d_now,
                              int32_t* d_est, uint8_t* d_drop, int32_t* d_order, int32_t* d_seg_ptr,
                              uint32_t* d_status, void* stream);

/*
 * Drop-mask stream compaction: the survivor queues that go on to batching (Section 4.1,
 * the Request Broker keeps or drops each request; kept requests form the next batches).
 *
 *   max_snapshot_requests  promised upper bound on the requests of one snapshot, as for
 *                          pard_estimate_drop: from 2049 to PARD_FUSED_SNAPSHOT_CAPACITY every
 *                          snapshot is compacted by one workgroup, below and above that the
 *                          queues are compacted as one stream (where the bound plays no
 *                          further role).  A snapshot larger than the workgroup chosen for
 *                          such a bound can hold (the bound rounded up to 4096 or 8192)
 *                          raises bit 0 of the status word; the outputs are then unspecified
 *                          (never out of bounds)
 *                          Neither form makes a workgroup wait for another one: like every call
 *                          here it may share the device with other work on other streams.
 *   d_order, d_seg_ptr     as written by pard_estimate_drop
 *   d_drop                 device uint8[n], request order; zero = keep, anything else = drop
 *   d_surv_idx             device out int32[n] (capacity): d_order with dropped requests
 *                          removed, same order; entries past surv_ptr[K*S] are untouched
 *   d_surv_ptr             device out int32[K*S+1] offsets of the survivor queues
 *
 * Errors: PARD_E_NULL, PARD_E_BAD_SHAPE (n < 0, n >= 2^30, negative bound),
 * PARD_E_WORKSPACE, PARD_E_HIP.
 */
int pard_compact(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                 const int32_t* d_order, const int32_t* d_seg_ptr, const uint8_t* d_drop,
                 int32_t* d_surv_idx, int32_t* d_surv_ptr,
                 void* d_workspace, int64_t workspace_bytes, void* stream);

/*
 * The whole path in one call: pard_estimate_drop followed by pard_compact, with the same outputs
 * (Section 3.2 Eq.(1),(2),(4) for the estimate, Section 3.3 for the order, Section 4.1 for the kept
 * requests that go on to batching).  Where the estimate kernels see a snapshot's queues complete in
 * on-chip memory (promised bounds from 2049 to PARD_FUSED_SNAPSHOT_CAPACITY) they also count and stage
 * its survivors, so that the compaction step neither counts nor reads d_order and d_drop again; for
 * every other shape the call is the two calls one after the other.
 *
 *   d_surv_idx, d_surv_ptr   as for pard_compact
 *   between_event            NULL, or a hipEvent_t that the call records on `stream` between the kernels of
 *                            the estimate step and those of the compaction step (lets a caller time the steps)
 *   everything else          as for pard_estimate_drop; the workspace must have the size pard_workspace_bytes
 *                            reports (it holds one staged survivor slot per request on top of what the two
 *                            separate calls need)
 * Errors: those of pard_estimate_drop and pard_compact.
 */
int pard_estimate_drop_compact(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                               const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                               const int32_t* d_snap_ptr, const int32_t* d_now,
                               int32_t* d_est, uint8_t* d_drop, int32_t* d_order, int32_t* d_seg_ptr,
                               int32_t* d_surv_idx, int32_t* d_surv_ptr,
                               void* d_workspace, int64_t workspace_bytes, void* between_event, void* stream);

/* Variants of the downstream latency (Section 5.1 baseline table; Section 5.3 ablations). */
enum { PARD_SUB_FULL = 0,        /* sum q_i + sum d_i + w, w = sampled lambda-quantile of the batch wait */
       PARD_SUB_LOWER = 1,       /* batch wait assumed 0            (the "-lower" ablation)                */
       PARD_SUB_UPPER = 2,       /* batch wait assumed sum d_i      (the "-upper" ablation)                */
       PARD_SUB_SF = 3,          /* sum d_i only: ignores Q and W of later modules ("-sf")                 */
       PARD_SUB_BACK = 4 };      /* 0: preceding and current modules only ("-back")                        */

#define PARD_MAX_WAIT_SAMPLES 16384        /* samples of the arrival process, at most                     */
#define PARD_MAX_WAIT_LATENCY (1 << 25)    /* the sampled variant needs every latency entry <= this       */

/*
 * Queue lengths: d_qlen[u*S + s] = number of requests of snapshot u whose (clamped) stage is
 * s - the monitored queue state the State Planner works from (Section 4.1, step 1).
 *
 *   d_stage, d_snap_ptr    device, as for pard_estimate_drop
 *   d_qlen                 device out int32[K*S]
 * Errors: PARD_E_NULL, PARD_E_BAD_SHAPE, PARD_E_HIP.  Enqueues on `stream`, allocates nothing.
 */
int pard_queue_lengths(const pard_plan_t* plan, int64_t n, const int32_t* d_stage, const int32_t* d_snap_ptr,
                       int32_t* d_qlen, void* stream);

/*
 * The State Planner's part of Eq.(4) (Section 3.2, "Batch wait estimation"): per (snapshot,
 * stage) the latency of the modules after it, maximum over the downstream DAG paths,
 *   L_sub = sum q_i + sum d_i + w
 * with q_i = floor(ceil(n_i/B_i) * lat_i[B_i] / W_i), d_i = lat_i[min(B_i, n_i + 1)], n_i = d_qlen,
 * and w the lambda-quantile (lambda = lambda_num / lambda_den) of the aggregated batch wait
 * time, sampled from the collected arrival process: sample j draws for every stage i the
 * arrival a = max(d_samples[d_picks[j*S + i] mod num_samples], 0), which waits
 * (d_i - a mod d_i) mod d_i for module i's next batch; the waits of a path's later stages add up
 * to T_j; w is the ceil(lambda * num_samples)-th smallest T_j (lambda = 0: 0, lambda = 1: sum d_i).
 * The random draws are the caller's (d_picks); nothing is generated here.
 *
 *   variant                PARD_SUB_*; only PARD_SUB_FULL reads lambda, samples and picks
 *   d_qlen                 device int32[K*S], >= 0 (negative values read as 0)
 *   num_samples            1..PARD_MAX_WAIT_SAMPLES (the paper's default is 10,000)
 *   d_samples              device int32[num_samples] arrival times, microseconds
 *   d_picks                device uint32[num_samples * S]
 *   d_sub                  device out int64[K*S], microseconds, saturated at 2^40
 * Errors: PARD_E_NULL, PARD_E_BAD_SHAPE (variant, lambda outside [0,1], sample count),
 * PARD_E_UNSUPPORTED (PARD_SUB_FULL with a latency entry above PARD_MAX_WAIT_LATENCY), PARD_E_HIP.
 * Enqueues on `stream`, allocates nothing; the sampled variant stages the drawn arrivals in
 * scratch memory the plan owns, so two such calls on one plan must not run at the same time.
 */
int pard_sub_latency(const pard_plan_t* plan, const int32_t* d_qlen, int32_t variant,
                     int64_t lambda_num, int64_t lambda_den, int32_t num_samples,
                     const int32_t* d_samples, const uint32_t* d_picks, int64_t* d_sub, void* stream);

/*
 * The monitored queueing delay q_i of every (snapshot, stage) (Section 3.2, State Planner: the
 * recent average queueing delay from a sliding window, by default 5 s and linearly weighted).
 * Series u*S + s holds series_len samples, in any order: a request left that queue at
 * d_time[(u*S + s)*series_len + j] after waiting d_delay[...] there (microseconds, negative
 * delays read as 0).  Seen from d_now[u], a sample of age = now - time weighs window_us - age
 * when 0 <= age < window_us and nothing otherwise (pad unused slots with a time after now);
 *   d_q[u*S + s] = floor(sum w * delay / sum w),  0 when no sample lies in the window.
 *
 *   series_len             0..PARD_MAX_DELAY_SAMPLES
 *   window_us              1..2^31-1
 *   d_time, d_delay        device int32[K*S*series_len]
 *   d_now                  device int32[K]
 *   d_q                    device out int32[K*S]
 * Errors: PARD_E_NULL, PARD_E_BAD_SHAPE, PARD_E_HIP.  Enqueues on `stream`, allocates nothing.
 */
#define PARD_MAX_DELAY_SAMPLES (1 << 30)
int pard_queue_delay(const pard_plan_t* plan, int32_t series_len, int64_t window_us, const int32_t* d_time,
                     const int32_t* d_delay, const int32_t* d_now, int32_t* d_q, void* stream);

/*
 * pard_sub_latency with the monitored queueing delays in place of the ones derived from the
 * queue lengths: q_i = max(d_qdelay[u*S + i], 0) (e.g. the output of pard_queue_delay); d_i still
 * follows d_qlen.  Everything else as for pard_sub_latency; d_qdelay NULL is PARD_E_NULL.
 */
int pard_sub_latency_q(const pard_plan_t* plan, const int32_t* d_qlen, const int32_t* d_qdelay, int32_t variant,
                       int64_t lambda_num, int64_t lambda_den, int32_t num_samples,
                       const int32_t* d_samples, const uint32_t* d_picks, int64_t* d_sub, void* stream);

/*
 * pard_estimate_drop with the downstream part given (Eq.(4): the Request Broker adds its own
 * stage's wait and execution to the State Planner's L_sub):
 *   est = cost_k(pos) + d_sub[u*S + k]      (d_sub >= 0; values above 2^40 read as 2^40)
 * Everything else as pard_estimate_drop.
 */
int pard_estimate_drop_sub(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                           const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                           const int32_t* d_snap_ptr, const int32_t* d_now, const int64_t* d_sub,
                           int32_t* d_est, uint8_t* d_drop, int32_t* d_order, int32_t* d_seg_ptr,
                           void* d_workspace, int64_t workspace_bytes, void* stream);

/*
 * Sequentially consistent dropping: the Request Broker takes the requests of a queue in queue
 * order and decides each one before the next (Section 4.1); a dropped request never takes a
 * batch slot, so the position that enters a request's own-stage cost is the number of requests
 * ahead of it in its queue that were KEPT, not all of them.  Everything else as
 * pard_estimate_drop (d_sub == NULL) or pard_estimate_drop_sub (d_sub given).  d_order and
 * d_seg_ptr are the same as in the one-pass calls; d_est and d_drop differ.  Both snapshot
 * sizes are served (on chip up to PARD_FUSED_SNAPSHOT_CAPACITY requests, after the sort above).
 */
int pard_estimate_drop_consistent(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                                  const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                                  const int32_t* d_snap_ptr, const int32_t* d_now, const int64_t* d_sub,
                                  int32_t* d_est, uint8_t* d_drop, int32_t* d_order, int32_t* d_seg_ptr,
                                  void* d_workspace, int64_t workspace_bytes, void* stream);

/*
 * Ranked downstream positions: pard_estimate_drop, except that in a later queue a request does
 * not join the back but takes the place its budget gives it.  The queues are kept in
 * remaining-budget order (Section 3.3), so at a later stage i the requests ahead of a newcomer
 * with deadline d are those that order serves first - deadline <= d under PARD_ORDER_LBF (the
 * requests already there win ties), deadline >= d under PARD_ORDER_HBF, the whole queue under
 * PARD_ORDER_FCFS - and
 *   est = cost_k(pos) + max over the paths through k of sum over later stages i of cost_i(ahead_i(d)).
 * d_order and d_seg_ptr are the same as in pard_estimate_drop; d_est and d_drop differ.
 * Arguments, workspace and errors as for pard_estimate_drop; both snapshot sizes are served.
 */
int pard_estimate_drop_ranked(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                              const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                              const int32_t* d_snap_ptr, const int32_t* d_now,
                              int32_t* d_est, uint8_t* d_drop, int32_t* d_order, int32_t* d_seg_ptr,
                              void* d_workspace, int64_t workspace_bytes, void* stream);

/*
 * Adaptive request priority with delayed transition (Section 3.3).  Per (snapshot u, stage s), from
 * the series d_rate[(u*S + s)*series_len + t] of the module's monitored input workload T_in
 * (requests per second, >= 0):
 *   T_m     = W * B * 10^6 / lat[B] requests per second        the module's throughput
 *   T_s[t]  = floor(mean of the last `window` samples up to t)  the sliding-window average
 *   eps     = sum |T_in - T_s| / sum T_in                       (0 for an all-zero series)
 *   mu[t]   = T_in[t] / T_m
 *   HBF when mu[t] > 1 + eps, LBF when mu[t] < 1 - eps, unchanged in between, starting from
 *   d_prev_mode[u*S + s] (PARD_ORDER_LBF when d_prev_mode is NULL).
 * d_mode[u*S + s] receives the priority in force after the last sample (PARD_ORDER_LBF or
 * PARD_ORDER_HBF).  All comparisons are exact (cross-multiplied integers).
 * Errors: PARD_E_NULL, PARD_E_BAD_SHAPE (series_len < 1, window < 1), PARD_E_HIP.
 */
int pard_priority_modes(const pard_plan_t* plan, int32_t series_len, int32_t window, const int32_t* d_rate,
                        const int32_t* d_prev_mode, int32_t* d_mode, void* stream);

/*
 * Installs queue orders in a plan: d_mode holds one PARD_ORDER_LBF / PARD_ORDER_HBF per stage
 * record (S entries for a plan with one shared DAG, K*S otherwise, e.g. the output of
 * pard_priority_modes).  The update is enqueued on `stream`; calls that use the plan must be
 * ordered after it, and no other stream may be using the plan meanwhile.  A stage that was
 * PARD_ORDER_FCFS loses that order.
 */
int pard_plan_set_modes(pard_plan_t* plan, const int32_t* d_mode, void* stream);

/*
 * Reactive dropping policies on the same snapshot (Section 5.1, "Baselines"): what the proactive estimate is
 * compared with.  Both write a drop mask in request order like pard_estimate_drop; neither looks at the modules
 * after the current one.
 *
 * PARD_REACTIVE_WINDOW_SCAN - the policy the paper describes for Nexus: every queue is scanned in the order
 *   given (d_order/d_seg_ptr as written by pard_estimate_drop; a plan whose stages use PARD_ORDER_FCFS gives
 *   the paper's arrival order) with a window of one batch.  With n requests in the queue the window at position
 *   p holds w = min(B, n - p) requests, runs as one batch of w and ends at now + lat[w]; it fits when no
 *   deadline in it is earlier.  d_first_kept[u*S + s] = the first position whose window fits (n when none
 *   does); the requests before it are dropped, all others kept.
 *     reads d_deadline, d_now, d_order, d_seg_ptr; d_arrival, d_stage, d_snap_ptr may be NULL
 * PARD_REACTIVE_SLO_SPLIT - Clipper++: the end-to-end SLO (deadline - arrival) is divided among the modules in
 *   proportion to their execution durations d_i = lat_i[B_i], SLO_k = SLO d_k / sum d_i; a request at module k
 *   is dropped once the time since it was sent exceeds the budgets of the modules up to and including k:
 *   now - arrival > SLO P_k / T_k (exactly, no rounding), P_k = summed durations along the longest way from a
 *   source to k, T_k = P_k + the longest way from k to a sink.  For one module this is Clipper's own rule,
 *   now > deadline; T_k = 0 reads as P_k / T_k = 1.
 *     reads d_arrival, d_deadline, d_stage, d_snap_ptr, d_now; d_order, d_seg_ptr, d_first_kept may be NULL
 *
 *   d_drop        device out uint8[n], 1 = drop, request order
 *   d_first_kept  device out int32[K*S] (window scan only)
 * Errors: PARD_E_NULL, PARD_E_BAD_SHAPE (policy, n), PARD_E_UNSUPPORTED (SLO split with a path whose summed
 * durations reach 2^30 microseconds), PARD_E_HIP.  Enqueues on `stream`, allocates nothing.
 */
enum { PARD_REACTIVE_WINDOW_SCAN = 0, PARD_REACTIVE_SLO_SPLIT = 1 };
int pard_reactive_drop(const pard_plan_t* plan, int32_t policy, int64_t n,
                       const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                       const int32_t* d_snap_ptr, const int32_t* d_now, const int32_t* d_order, const int32_t* d_seg_ptr,
                       uint8_t* d_drop, int32_t* d_first_kept, void* stream);

/* Static, human-readable text for a status code. */
const char* pard_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* PARD_H_ */
